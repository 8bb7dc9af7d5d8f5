// Host-thread executor behind tests/cpu_emul/hip/hip_runtime.h (test infrastructure only).
#include <hip/hip_runtime.h>

namespace hip_emul {
thread_local dim3 t_threadIdx, t_blockIdx;
dim3 g_blockDim, g_gridDim;
thread_local Wave* t_wave = nullptr;
pthread_barrier_t g_block_bar;
alignas(16) float g_dynamic_lds[40960];  // 160 KB, the LDS of one CU

void launch(dim3 grid, dim3 block, void (*body)(void*), void* closure) {
  const unsigned nthreads = block.x * block.y * block.z;
  const unsigned nwaves = (nthreads + 63) / 64;
  if (nthreads % 64 != 0) {
    fprintf(stderr, "hip_emul: block size %u is not a multiple of the wavefront size\n", nthreads);
    abort();
  }
  g_blockDim = block;
  g_gridDim = grid;
  std::vector<Wave> waves(nwaves);
  for (auto& w : waves) pthread_barrier_init(&w.bar, nullptr, 64);
  pthread_barrier_init(&g_block_bar, nullptr, nthreads);
  pthread_barrier_t between;
  pthread_barrier_init(&between, nullptr, nthreads);
  std::vector<std::thread> pool;
  pool.reserve(nthreads);
  for (unsigned tid = 0; tid < nthreads; ++tid) {
    pool.emplace_back([&, tid] {
      t_threadIdx = dim3(tid % block.x, (tid / block.x) % block.y, tid / (block.x * block.y));
      t_wave = &waves[tid / 64];
      for (unsigned bz = 0; bz < grid.z; ++bz)
        for (unsigned by = 0; by < grid.y; ++by)
          for (unsigned bx = 0; bx < grid.x; ++bx) {
            t_blockIdx = dim3(bx, by, bz);
            body(closure);
            pthread_barrier_wait(&between);  // workgroups run one after the other
          }
    });
  }
  for (auto& th : pool) th.join();
  for (auto& w : waves) pthread_barrier_destroy(&w.bar);
  pthread_barrier_destroy(&g_block_bar);
  pthread_barrier_destroy(&between);
}
}  // namespace hip_emul

