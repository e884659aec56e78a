// TEST INFRASTRUCTURE: the batching server (csrc/batcher.cpp) compiled by g++ under
// ThreadSanitizer against the CPU stand-in for HIP, with the preprocessing handle replaced by
// a stub that only records what it is given.  It checks the server's own threading: several
// threads submit, several collect, every request must come back exactly once, in a batch no
// larger than batch_max, carrying its own bytes.  No GPU, no kernels.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/prep.h"

// ---- stub of the handle API that the server calls -----------------------------------------
struct prep_handle {
    int32_t max_batch;
    std::vector<int32_t> status;
};

extern "C" {

int prep_create(prep_handle **out, const prep_config *cfg)
{
    *out = new prep_handle{cfg->max_batch, {}};
    return PREP_OK;
}

int prep_destroy(prep_handle *h)
{
    delete h;
    return PREP_OK;
}

// "Decodes" a batch: the slab of image i gets the first bytes of its file (a tag the driver
// put there); a file that starts with 'X' is reported corrupt.
int prep_decode_resize_batch(prep_handle *h, const uint8_t *bits, const uint64_t *offsets, int32_t n,
                             const prep_params *params, void *out, void *)
{
    if (n > h->max_batch) return PREP_E_TOO_LARGE;
    const size_t slab = (size_t)3 * params->crop_h * params->crop_w * sizeof(float);
    h->status.assign((size_t)n, PREP_OK);
    for (int32_t i = 0; i < n; i++) {
        const uint8_t *f = bits + offsets[i];
        const size_t len = (size_t)(offsets[i + 1] - offsets[i]);
        if (f[0] == 'X') h->status[(size_t)i] = PREP_E_CORRUPT;
        memset((uint8_t *)out + (size_t)i * slab, 0, slab);
        memcpy((uint8_t *)out + (size_t)i * slab, f, len < slab ? len : slab);
    }
    std::this_thread::sleep_for(std::chrono::microseconds(150 + 20 * n));  // the "GPU" at work
    return PREP_OK;
}

int prep_get_status(prep_handle *h, int32_t *status, int32_t n)
{
    for (int32_t i = 0; i < n; i++) status[i] = h->status[(size_t)i];
    return PREP_OK;
}

}  // extern "C"

// ---- driver --------------------------------------------------------------------------------
int main(int argc, char **argv)
{
    const int n_submitters = argc > 1 ? atoi(argv[1]) : 4;
    const int per_submitter = argc > 2 ? atoi(argv[2]) : 500;
    const int n_collectors = 2;
    const int total = n_submitters * per_submitter;
    prep_server_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.handle.device = 0;
    cfg.handle.max_width = cfg.handle.max_height = 16;
    cfg.handle.max_bitstream_bytes = 1;
    cfg.params.crop_h = cfg.params.crop_w = 2;
    cfg.params.out_dtype = PREP_F32;
    cfg.params.filter = PREP_FILTER_BILINEAR;
    cfg.n_consumers = 3;
    cfg.batch_max = 8;
    cfg.time_queue_us = 300;
    cfg.max_request_bytes = 64;
    cfg.queue_capacity = 64;
    prep_server *s = nullptr;
    if (prep_server_create(&s, &cfg) != PREP_OK) { fprintf(stderr, "create failed\n"); return 2; }

    std::vector<std::atomic<int>> seen((size_t)total);
    for (auto &x : seen) x = 0;
    std::atomic<int> collected{0}, refused{0}, wrong{0};
    std::vector<std::thread> threads;
    for (int c = 0; c < n_collectors; c++)
        threads.emplace_back([&] {
            while (collected.load() < total) {
                prep_server_result r;
                const int got = prep_server_next(s, &r, 20000);
                if (got != 1) continue;
                uint8_t slab[48];
                if (prep_server_copy_tensor(s, &r, slab) != PREP_OK) wrong++;
                uint64_t tag;
                memcpy(&tag, slab + 1, 8);
                const bool corrupt = slab[0] == 'X';
                if (tag != r.tag || r.batch_size < 1 || r.batch_size > cfg.batch_max || r.consumer < 0 ||
                    r.consumer >= cfg.n_consumers || r.arrival_ns > r.start_ns || r.start_ns > r.done_ns ||
                    r.status != (corrupt ? PREP_E_CORRUPT : PREP_OK) || r.tag >= (uint64_t)total)
                    wrong++;
                else
                    seen[(size_t)r.tag]++;
                if (prep_server_release(s, &r) != PREP_OK) wrong++;
                collected++;
            }
        });
    for (int t = 0; t < n_submitters; t++)
        threads.emplace_back([&, t] {
            for (int k = 0; k < per_submitter; k++) {
                const uint64_t tag = (uint64_t)t * per_submitter + k;
                uint8_t file[24];
                memset(file, 0, sizeof file);
                file[0] = tag % 17 == 3 ? 'X' : 'J';
                memcpy(file + 1, &tag, 8);
                // the queue is small on purpose: a refused request is offered again
                while (prep_server_submit(s, file, 9 + tag % 15, tag) != PREP_OK) {
                    refused++;
                    std::this_thread::sleep_for(std::chrono::microseconds(50));
                }
                if (k % 64 == 63) std::this_thread::sleep_for(std::chrono::microseconds(400));  // idle gaps
            }
        });
    for (auto &th : threads) th.join();
    int bad = wrong.load();
    for (auto &x : seen) bad += x.load() != 1;
    prep_server_result r;
    if (prep_server_next(s, &r, 1000) != 0) bad++;  // nothing is left
    prep_server_destroy(s);
    printf("requests %d refused-and-retried %d bad %d\n", total, refused.load(), bad);
    return bad ? 1 : 0;
}
