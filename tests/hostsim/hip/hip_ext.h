#pragma once
#define hipExtLaunchKernelGGL(kernel, grid, block, shmem, stream, e0, e1, flags, ...) hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__)
