#include <hip/hip_runtime.h>
#include <thread>
#include <vector>
#include <string>

namespace emu {
thread_local dim3 t_threadIdx, t_blockIdx, t_blockDim, t_gridDim;
thread_local Block* t_block;

// EMU_BLOCKS: "all", or a stride N (every N-th block plus the last), default 1 = all
void launch(unsigned grid, unsigned block, size_t lds, const std::function<void()>& body)
{
    // EMU_BLOCKS: comma list of block ranges "a-b" or single blocks to run (default: all)
    const char* env = getenv("EMU_BLOCKS");
    std::vector<std::pair<unsigned, unsigned>> ranges;
    if (env && *env) {
        std::string s(env);
        size_t pos = 0;
        while (pos < s.size()) {
            size_t q = s.find(',', pos);
            if (q == std::string::npos) q = s.size();
            std::string item = s.substr(pos, q - pos);
            size_t dash = item.find('-');
            unsigned a = (unsigned)atoi(item.c_str());
            unsigned e = dash == std::string::npos ? a : (unsigned)atoi(item.c_str() + dash + 1);
            ranges.push_back({a, e});
            pos = q + 1;
        }
    }
    for (unsigned b = 0; b < grid; ++b) {
        bool run = ranges.empty();
        for (auto& r : ranges) run = run || (b >= r.first && b <= r.second);
        if (!run) continue;
        if (getenv("EMU_VERBOSE")) { fprintf(stderr, "[emu] block %u of %u (%u threads, %zu B LDS)\n", b, grid, block, lds); }
        Block blk;
        blk.nthreads = (int)block;
        blk.lds_bytes = lds;
        blk.lds = (unsigned char*)malloc(lds ? lds : 1);           // exact size: ASan sees LDS overruns
        memset(blk.lds, 0xA5, lds);
        pthread_barrier_init(&blk.all, nullptr, block);
        const unsigned nwaves = (block + 63) / 64;
        for (unsigned w = 0; w < nwaves; ++w)
            pthread_barrier_init(&blk.wave[w], nullptr, std::min(64u, block - w * 64));
        for (unsigned h = 0; h < (block + 31) / 32; ++h)
            pthread_barrier_init(&blk.half[h], nullptr, std::min(32u, block - h * 32));
        std::vector<std::thread> th;
        th.reserve(block);
        for (unsigned t = 0; t < block; ++t)
            th.emplace_back([&, t]() {
                t_threadIdx = dim3(t); t_blockIdx = dim3(b); t_blockDim = dim3(block); t_gridDim = dim3(grid);
                t_block = &blk;
                body();
            });
        for (auto& x : th) x.join();
        for (unsigned w = 0; w < nwaves; ++w) pthread_barrier_destroy(&blk.wave[w]);
        for (unsigned h = 0; h < (block + 31) / 32; ++h) pthread_barrier_destroy(&blk.half[h]);
        pthread_barrier_destroy(&blk.all);
        free(blk.lds);
    }
}
}  // namespace emu
