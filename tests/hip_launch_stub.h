/*
 * Test-only: force-included (-include) ahead of the library's sources when they are built for the
 * HOST with AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_host_sanitizers.py).
 * Every HIP call the host code makes succeeds and does nothing, so that the planning,
 * validation and launch-shape code of every entry point runs to its end on a machine without
 * a GPU, on device pointers that are never dereferenced.  The real header is included first;
 * its include guard keeps the sources' own #include from undoing the replacements.
 */
#include <hip/hip_runtime.h>
#include <string.h>

#undef hipLaunchKernelGGL
#define hipLaunchKernelGGL(kernel, grid, block, lds, stream, ...) adaptra_stub_launch((grid), (block), (size_t)(lds))
static inline void adaptra_stub_launch(dim3 grid, dim3 block, size_t lds) {
    /* what a real launch would refuse */
    if (grid.x < 1 || grid.x > 2147483647u || block.x < 1 || block.x > 1024 || lds > 160 * 1024) __builtin_trap();
}
#define hipGetLastError() hipSuccess
#define hipFuncSetAttribute(...) hipSuccess
#define hipStreamSynchronize(stream) hipSuccess
#define hipEventRecord(event, stream) hipSuccess
#define hipMemcpyAsync(dst, src, bytes, kind, stream) \
    ((kind) == hipMemcpyDeviceToHost ? (memset((dst), 0, (bytes)), hipSuccess) : hipSuccess)
#define hipGetDevice(out) (*(out) = 0, hipSuccess)
#define hipGetSymbolAddress(out, symbol) (*(out) = (void *)(uintptr_t)0x100000, hipSuccess)
