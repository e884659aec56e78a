// Lane scheduler of the CPU stand-in for HIP (test infrastructure).
#include <hip/hip_runtime.h>

namespace hip_emul {

void launch(dim3 grid, dim3 block, const std::function<void()> &fn)
{
    const unsigned n = block.x * block.y * block.z;
    for (unsigned bz = 0; bz < grid.z; bz++)
        for (unsigned by = 0; by < grid.y; by++)
            for (unsigned bx = 0; bx < grid.x; bx++) {
                BlockCtx ctx(n);
                std::vector<std::thread> lanes;
                lanes.reserve(n);
                for (unsigned t = 0; t < n; t++)
                    lanes.emplace_back([&, t]() {
                        ThreadState &s = tls;
                        s.tid = dim3(t % block.x, (t / block.x) % block.y, t / (block.x * block.y));
                        s.bid = dim3(bx, by, bz);
                        s.bdim = block;
                        s.gdim = grid;
                        s.ctx = &ctx;
                        s.or_calls = 0;
                        fn();
                        // a lane that has returned no longer takes part in barriers
                        ctx.wave_bar[t >> 6]->arrive_and_drop();
                        ctx.bar.arrive_and_drop();
                    });
                for (auto &l : lanes) l.join();
            }
}

}  // namespace hip_emul
