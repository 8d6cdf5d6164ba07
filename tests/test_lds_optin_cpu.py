"""Host-side bookkeeping of the large-LDS opt-in (csrc/lds_optin.h): the opt-in is remembered per kernel
function address and device, so two kernel instantiations that share a function-pointer TYPE (every
instantiation of one template does) are each reported as needing their own attribute call.  The header has
no GPU dependency; this compiles a small program against it with the host compiler."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r'''
#include <cstdio>
#include "lds_optin.h"
template <int V> void kernel_like(int*, float) {}      // two instantiations, one pointer type
template <class KernelT> int calls_needed(KernelT k, int dev) {      // mirrors allow_lds(): generic over the pointer type
  auto& reg = aa::lds_optin_registry();
  if (!reg.needs((const void*)k, dev)) return 0;
  reg.done((const void*)k, dev);      // stands for a successful hipFuncSetAttribute
  return 1;
}
int main() {
  int n = 0;
  n += calls_needed(kernel_like<0>, 0);      // 1: first sight of this function on device 0
  n += calls_needed(kernel_like<1>, 0);      // 1: same pointer type, other function
  n += calls_needed(kernel_like<0>, 0);      // 0: already done
  n += calls_needed(kernel_like<0>, 1);      // 1: other device
  n += calls_needed(kernel_like<1>, 0);      // 0
  std::printf("%d %zu\n", n, aa::lds_optin_registry().size());
  return 0;
}
'''


def test_optin_is_keyed_by_function_and_device(tmp_path):
    src = tmp_path / "optin.cpp"
    exe = tmp_path / "optin"
    src.write_text(PROGRAM)
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", os.path.join(ROOT, "paper_2312_08874_amd", "csrc"), "-o", str(exe),
                    str(src), "-lpthread"], check=True)
    out = subprocess.run([str(exe)], check=True, stdout=subprocess.PIPE).stdout.decode().split()
    assert out == ["3", "3"], out
