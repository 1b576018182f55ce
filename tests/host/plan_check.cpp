// The library's host-side planning and argument validation (paper_2501_16007_amd/csrc/plan.hpp, the
// very header the HIP library compiles) built for the host alone with the address and
// undefined-behaviour sanitizers, and driven without a GPU: the rejection cases of the C ABI, and
// the invariants every plan must keep (parts cover the chunk, slot ranges of segments never overlap
// and stay inside the launch, sizes do not overflow) over a sweep of sizes including the extremes.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <vector>

#include "../../paper_2501_16007_amd/csrc/plan.hpp"

using namespace toploc::plan;

static int failures = 0;
#define CHECK(cond)                                                             \
    do {                                                                        \
        if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++failures; } \
    } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd()
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return rng_state;
}

static void check_parameters()
{
    toploc_params ok = {128, 32, 4096, TOPLOC_PRIME};
    CHECK(chunk_len(&ok) == 131072);
    CHECK(chunk_len(nullptr) == 0);
    toploc_params p = ok;
    p.k = 0; CHECK(chunk_len(&p) == 0);
    p = ok; p.k = TOPLOC_MAX_K + 1; CHECK(chunk_len(&p) == 0);
    p = ok; p.k = TOPLOC_MAX_K_TOPK; CHECK(chunk_len(&p, TOPLOC_MAX_K_TOPK) == 131072);
    p = ok; p.prime = 65521; CHECK(chunk_len(&p) == 0);
    p = ok; p.hidden = 3; CHECK(chunk_len(&p) == 0);              // N = 96 < k
    p = ok; p.chunk_tokens = 3; p.hidden = 5; p.k = 8; CHECK(chunk_len(&p) == 0);   // N % 8 != 0
    p = ok; p.chunk_tokens = 1u << 16; p.hidden = 1u << 16; CHECK(chunk_len(&p) == 0);   // N = 2^32
    p = ok; p.chunk_tokens = 0; CHECK(chunk_len(&p) == 0);
    p = ok; p.chunk_tokens = 0xFFFFFFFFu; p.hidden = 0xFFFFFFF8u; CHECK(chunk_len(&p) == 0);   // no overflow on the way
    toploc_params f = {128, 32, 4096, TOPLOC_PRIME32};
    CHECK(chunk_len_mixed(&f, TOPLOC_DTYPE_F32, TOPLOC_DTYPE_F32) == 131072);
    CHECK(chunk_len_mixed(&f, TOPLOC_DTYPE_BF16, TOPLOC_DTYPE_BF16) == 0);    // the prime follows the proof's precision
    CHECK(chunk_len_mixed(&ok, TOPLOC_DTYPE_F32, TOPLOC_DTYPE_BF16) == 131072);
    CHECK(chunk_len_mixed(&ok, 2, TOPLOC_DTYPE_BF16) == 0);
    f.k = TOPLOC_MAX_K_F32 + 1; CHECK(chunk_len_mixed(&f, TOPLOC_DTYPE_F32, TOPLOC_DTYPE_F32) == 0);
}

static void check_rejections()
{
    const void* fake = (const void*)(uintptr_t)0x10000;      // never dereferenced
    const void* odd = (const void*)(uintptr_t)0x10001;
    const void* mis8 = (const void*)(uintptr_t)0x10008;
    const uint64_t n = 131072;
    CHECK(check_fixed(n, 1, fake, fake, 2, fake, 1, fake) == kGo);
    CHECK(check_fixed(0, 1, fake, fake, 2, fake, 1, fake) == TOPLOC_EINVAL);
    CHECK(check_fixed(n, 1ull << 31, fake, fake, 2, fake, 1, fake) == TOPLOC_EINVAL);
    CHECK(check_fixed(n, 0, nullptr, nullptr, 2, nullptr, 1, nullptr) == TOPLOC_OK);       // empty batch: nothing is looked at
    CHECK(check_fixed(n, 1, nullptr, fake, 2, fake, 1, fake) == TOPLOC_EINVAL);
    CHECK(check_fixed(n, 1, mis8, fake, 2, fake, 1, fake) == TOPLOC_EINVAL);
    CHECK(check_fixed(n, 1, fake, odd, 2, fake, 1, fake) == TOPLOC_EINVAL);
    CHECK(check_fixed(n, 1, fake, fake, 2, odd, 4, fake) == TOPLOC_EINVAL);
    CHECK(check_fixed(n, 1, fake, fake, 2, odd, 1, fake) == kGo);
    CHECK(check_fixed(n, 1, fake, fake, 2, fake, 1, mis8) == TOPLOC_EINVAL);
    CHECK(check_fixed(n, 1, fake, fake, 2, fake, 1, nullptr) == kGo);                      // the workspace is optional
    // the library's fixed scratch
    const size_t scratch = TOPLOC_STATIC_SCRATCH_BYTES;
    CHECK(check_static_scratch(plan_fixed(16384, 32768, 0), 16384, 128, scratch) == kGo);       // fused
    CHECK(check_static_scratch(plan_fixed(16384, 32768, 0), 16384, 512, scratch) == TOPLOC_ESCRATCH);
    CHECK(check_static_scratch(plan_fixed(48, 16384, 0), 48, 512, scratch) == kGo);
    CHECK(check_static_scratch(plan_fixed(1000, 16384, 4096), 1000, 128, scratch) == TOPLOC_ESCRATCH);   // forced cut
    // segments
    SegmentPlan pl = plan_segments(2, 9, 4096, 128, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0);
    CHECK(pl.ok);
    const uint64_t* off = (const uint64_t*)fake;
    const size_t need = segments_workspace_bytes(pl, 128, 2);
    CHECK(check_segments(pl, 2, 128, TOPLOC_DTYPE_BF16, fake, off, fake, fake, 1, fake, need) == kGo);
    CHECK(check_segments(pl, 2, 128, TOPLOC_DTYPE_BF16, fake, off, fake, fake, 1, fake, need - 1) == TOPLOC_EWORKSPACE);
    CHECK(check_segments(pl, 2, 128, TOPLOC_DTYPE_F32, fake, off, fake, fake, 1, fake, need) == TOPLOC_EWORKSPACE);
    CHECK(check_segments(pl, 0, 128, TOPLOC_DTYPE_BF16, nullptr, nullptr, nullptr, nullptr, 1, nullptr, 0) == TOPLOC_OK);
    CHECK(check_segments(pl, 2, 128, TOPLOC_DTYPE_BF16, fake, nullptr, fake, fake, 1, fake, need) == TOPLOC_EINVAL);
    CHECK(check_segments(pl, 2, 128, TOPLOC_DTYPE_BF16, fake, (const uint64_t*)(uintptr_t)0x10004, fake, fake, 1, fake, need) ==
          TOPLOC_EINVAL);
    CHECK(check_segments(pl, 2, 128, TOPLOC_DTYPE_BF16, fake, off, fake, odd, 4, fake, need) == TOPLOC_EINVAL);
    CHECK(check_segments(pl, 2, 128, TOPLOC_DTYPE_BF16, fake, off, fake, fake, 1, nullptr, need) == TOPLOC_EINVAL);
    CHECK(!plan_segments(2, 9, 4100, 128, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0).ok);
    CHECK(!plan_segments(2, 9, 4096, 0, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0).ok);
    CHECK(!plan_segments(2, 9, 4096, 513, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0).ok);
    CHECK(!plan_segments(1ull << 31, 9, 4096, 128, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0).ok);
    CHECK(!plan_segments(2, ~0ull, 4096, 128, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0).ok);
    CHECK(!plan_segments(2, 9, 4096, 128, 5, TOPLOC_MAX_K, 0).ok);
    // running top-k, ring
    CHECK(stream_stride(128) == 16 + 512 + 256 && stream_stride(5) == 16 + 32 + 16);
    CHECK(stream_stride(128, TOPLOC_DTYPE_F32) == 16 + 512 + 512 && stream_stride(5, TOPLOC_DTYPE_F32) == 16 + 32 + 32);
    CHECK(stream_k_ok(512, TOPLOC_DTYPE_F32) && !stream_k_ok(513, TOPLOC_DTYPE_F32) && !stream_k_ok(128, 2) && !stream_k_ok(0));
    // one row per sequence
    CHECK(check_stream_append(fake, 4, fake, nullptr, nullptr, 4, 4096, 32, 0, 128) == kGo);
    CHECK(check_stream_append(fake, 4, fake, nullptr, nullptr, 4, 4096, 32, 32, 128) == TOPLOC_EINVAL);      // token >= chunk_tokens
    CHECK(check_stream_append(fake, 4, fake, nullptr, nullptr, 4, 4100, 32, 0, 128) == TOPLOC_EINVAL);
    CHECK(check_stream_append(fake, 4, fake, nullptr, nullptr, 4, 1u << 20, 1u << 12, 0, 128) == TOPLOC_EINVAL);
    CHECK(check_stream_append(nullptr, 4, fake, nullptr, nullptr, 4, 4096, 32, 0, 128) == TOPLOC_EINVAL);
    CHECK(check_stream_append(nullptr, 0, nullptr, nullptr, nullptr, 0, 4096, 32, 0, 128) == TOPLOC_OK);
    CHECK(check_stream_append(fake, 4, fake, nullptr, nullptr, 4, 4096, 32, 0, 513) == TOPLOC_EINVAL);
    CHECK(check_stream_append(fake, 4, fake, nullptr, nullptr, 4, 4096, 32, 0, 512, TOPLOC_DTYPE_F32) == kGo);
    CHECK(check_stream_append(fake, 4, fake, nullptr, nullptr, 4, 4096, 32, 0, 128, 7) == TOPLOC_EINVAL);
    // rows of any subset of the sequences
    CHECK(check_stream_append(fake, 8, fake, fake, fake, 3, 4096, 32, 99, 128) == kGo);                       // `token` is ignored
    CHECK(check_stream_append(fake, 0, fake, fake, fake, 3, 4096, 32, 0, 128) == TOPLOC_EINVAL);
    CHECK(check_stream_append(fake, 8, fake, fake, nullptr, 3, 4096, 32, 0, 128) == TOPLOC_EINVAL);
    CHECK(check_stream_append(fake, 8, fake, (const void*)(uintptr_t)0x10002, fake, 3, 4096, 32, 0, 128) == TOPLOC_EINVAL);
    CHECK(check_stream_append(fake, 8, fake, fake, fake, 0, 4096, 32, 0, 128) == TOPLOC_OK);
    CHECK(check_stream_emit(fake, 2, 128, fake, fake, false, nullptr, 0) == kGo);
    CHECK(check_stream_emit(fake, 2, 0, fake, fake, false, nullptr, 0) == TOPLOC_EINVAL);
    CHECK(check_stream_emit(fake, 2, 128, odd, fake, false, nullptr, 0) == TOPLOC_EINVAL);
    CHECK(check_stream_emit(fake, 2, 128, fake, fake, true, nullptr, 8) == TOPLOC_EINVAL);
    CHECK(check_stream_emit(fake, 0, 128, nullptr, nullptr, true, nullptr, 0) == TOPLOC_OK);
    CHECK(check_ring_append(fake, fake, 4, 12, 32) == TOPLOC_EINVAL);
    CHECK(check_ring_append(nullptr, nullptr, 0, 16, 32) == TOPLOC_OK);
    CHECK(check_ring_append(fake, mis8, 4, 16, 32) == TOPLOC_EINVAL);
}

// every fixed plan covers the chunk with whole parts, none of them empty except by a forced cut
static void check_fixed_plans()
{
    const uint64_t nvecs[] = {1, 2, 7, 1024, 4095, 4096, 4097, 16384, 20480, 32768, 65536, 65537, (1ull << 29) - 1};
    const uint64_t chunks[] = {1, 2, 3, 5, 64, 1000, 1023, 1024, 4096, 16384, (1ull << 31) - 1};
    const uint64_t forced[] = {0, 1, 2, 3, 7, 16, 4096};
    for (uint64_t nvec : nvecs)
        for (uint64_t nc : chunks)
            for (uint64_t fo : forced) {
                const FixedPlan f = plan_fixed(nc, nvec, fo);
                CHECK(f.parts >= 1 && f.part_vecs >= 1 && f.part_vecs <= nvec);
                CHECK((uint64_t)f.parts * f.part_vecs >= nvec);
                if (!fo) {
                    CHECK((uint64_t)(f.parts - 1) * f.part_vecs < nvec);          // the last part is not empty
                    CHECK(f.parts == 1 || (f.part_vecs >= kMinPartVecs && f.part_vecs % kRoundVecs == 0));
                    CHECK(f.part_vecs <= kMaxPartVecs || f.parts == 1);
                    if (nc >= kTargetGroups && nvec <= kMaxPartVecs) CHECK(f.parts == 1);
                }
                CHECK(cand_bytes(nc * f.parts, 512) >= nc * f.parts * 512 * 6);
            }
}

// Segments: with row offsets a_0 <= a_1 <= ... the slot ranges [a_i / pv + i, + ceil(len_i / pv)) are disjoint,
// ascending and inside the launch, whatever the lengths
static void check_segment_plans()
{
    for (int trial = 0; trial < 4000; ++trial) {
        const uint32_t hidden = 8u * (uint32_t)(1 + rnd() % 1024);
        const uint32_t dtype = (uint32_t)(rnd() % 2);
        const uint64_t n_seg = 1 + rnd() % 40;
        std::vector<uint64_t> off(n_seg + 1);
        uint64_t r = rnd() % 5;
        for (uint64_t i = 0; i <= n_seg; ++i) {
            off[i] = r;
            const uint64_t kind = rnd() % 6;
            r += kind == 0 ? 0 : kind == 1 ? 1 : kind == 2 ? 32 : kind == 3 ? rnd() % 100 : kind == 4 ? rnd() % 3000 : 2;
        }
        const uint64_t total_rows = off[n_seg] + rnd() % 3;
        const uint64_t forced = (rnd() % 3 == 0) ? 1 + rnd() % 9 : 0;
        const SegmentPlan pl = plan_segments(n_seg, total_rows, hidden, 128, dtype, TOPLOC_MAX_K_F32, forced);
        CHECK(pl.ok);
        if (!pl.ok) continue;
        CHECK(pl.row_vecs == hidden / (dtype ? 4 : 8) && pl.part_vecs >= 1 && pl.part_vecs <= kMaxSegmentVecs);
        uint64_t next_free = 0;
        for (uint64_t i = 0; i < n_seg; ++i) {
            const uint64_t a = off[i] * pl.row_vecs, len = (off[i + 1] - off[i]) * pl.row_vecs;
            const uint64_t first = a / pl.part_vecs + i, parts = (len + pl.part_vecs - 1) / pl.part_vecs;
            CHECK(first >= next_free);                  // no overlap with the segments before
            CHECK(first + parts <= pl.slots);           // inside the launch
            next_free = first + parts;
        }
        CHECK(segments_workspace_bytes(pl, 128, dtype ? 4 : 2) >= pl.slots * (128 * (dtype ? 8 : 6) + kPartDescBytes));
    }
    // the extremes: the most rows the plan accepts, one segment or very many
    const SegmentPlan big = plan_segments((1ull << 31) - 1, (1ull << 62) / 8, 8, 1, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0);
    CHECK(!big.ok || big.slots < (1ull << 31));
    const SegmentPlan one = plan_segments(1, 1ull << 20, 8192, 512, TOPLOC_DTYPE_BF16, TOPLOC_MAX_K, 0);
    CHECK(one.ok && one.part_vecs == kMaxPartVecs);
}

int main()
{
    check_parameters();
    check_rejections();
    check_fixed_plans();
    check_segment_plans();
    if (failures) { printf("%d check(s) failed\n", failures); return 1; }
    printf("plan_check ok\n");
    return 0;
}
