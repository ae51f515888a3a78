// Self-test of the wavefront primitives: each is compared, on the device, with a
// serial evaluation of its definition by lane 0.  Every access is to a fixed
// LDS array of 256 or 832 entries, so the test cannot touch memory it does not own.
#pragma once
#include "wave_ops.hpp"
#include "../../include/vms_replay.h"

__global__ __launch_bounds__(64) void selftest_kernel(u32 *fail)
{
    __shared__ u32 in[64], out[64];
    __shared__ u64 arr[256];
    __shared__ u64 big[832];
    __shared__ __attribute__((aligned(16))) uint16_t nar[2048];
    __shared__ __attribute__((aligned(16))) u32 nar32[2048];
    const u32 lane = lane_id();
    u32 bad = 0;
    for (u32 round = 0; round < 8; round++) {
        u32 v = (lane * 2654435761u + round * 40503u) ^ (lane << (round & 7));
        v = round == 7 ? 5u : (v >> (round * 3));
        in[lane] = v;
        wave_sync();
        // minimum
        u32 m = wave_min_u32(v), ref = 0xFFFFFFFFu;
        for (int i = 0; i < 64; i++) ref = min(ref, in[i]);
        if (m != ref) bad |= 1;
        // inclusive scan
        u32 tot, s = wave_scan_add(v & 0xFFFF, &tot);
        out[lane] = s;
        wave_sync();
        u32 run = 0;
        for (int i = 0; i < 64; i++) {
            run += in[i] & 0xFFFF;
            if (out[i] != run) bad |= 2;
        }
        if (tot != run) bad |= 4;
        // ballot / rank / lane reads
        u64 b = ballot((v & 1) != 0);
        u32 below = 0;
        for (u32 i = 0; i < lane; i++) below += in[i] & 1;
        if (rank_in(b) != below) bad |= 8;
        if (from_lane(v, (round * 9) & 63) != in[(round * 9) & 63]) bad |= 16;
        wave_sync();
    }
    // sorted-array helpers on a descending array of 150 keys, followed by zero keys as they require
    for (u32 i = lane; i < 256; i += 64) arr[i] = i < 150 ? (u64)(1000 - 3 * i) << 32 : 0;
    wave_sync();
    if (count_gt(arr, 150, (u64)700 << 32) != 100) bad |= 32;     // 1000-3i > 700  <=>  i < 100
    u32 c1, c2;
    count_gt2(arr, 150, ((u64)700 << 32) | 0xFFFFFFFFu, ((u64)700 << 32) - 1, &c1, &c2);
    if (c1 != 100 || c2 != 101) bad |= 32;
    for (u32 n = 1; n <= 150; n += (n < 70 ? 1 : 7)) {
        for (u32 i = lane; i < 256; i += 64) arr[i] = i < n ? (u64)(1000 - 3 * i) << 32 : 0;
        wave_sync();
        for (u32 probe = 540; probe <= 1003; probe += 1) {
            u64 key = ((u64)probe << 32) - 1;
            u32 ref = count_gt(arr, n, key), r = rank_desc(arr, n, key), r1, r2;
            rank_desc2(arr, n, key + ((u64)2 << 32), key, &r1, &r2);
            if (r != ref || r2 != ref || r1 != count_gt(arr, n, key + ((u64)2 << 32))) bad |= 256;
        }
        // the same ranks with the first search level cached in registers
        Probe pr;
        probe_refresh(pr, arr, n);
        for (u32 probe = 540; probe <= 1003; probe += 1) {
            u64 key = ((u64)probe << 32) - 1;
            if (rank_probe(pr, arr, n, key) != count_gt(arr, n, key)) bad |= 512;
        }
    }
    for (u32 i = lane; i < 256; i += 64) arr[i] = i < 150 ? (u64)(1000 - 3 * i) << 32 : 0;
    wave_sync();
    shift_up(arr, 70, 150);
    st_one(arr, 70u, (u64)12345);
    wave_sync();
    for (u32 i = 0; i < 151; i++) {
        u64 want = i < 70 ? (u64)(1000 - 3 * i) << 32 : (i == 70 ? (u64)12345 : (u64)(1000 - 3 * (i - 1)) << 32);
        if (arr[i] != want) bad |= 64;
    }
    shift_down(arr, 70, 151);
    for (u32 i = 0; i < 150; i++)
        if (arr[i] != (u64)(1000 - 3 * i) << 32) bad |= 128;
    for (u32 i = 151; i < 256; i++)
        if (arr[i] != 0) bad |= 128;                // the spare places stay zero (arr[150] keeps the moved key's copy)
    // the same over many tiles: 700 keys, 64 spare places, moved from places 0, 37 and 699
    for (u32 pos = 0; pos < 700; pos = pos == 0 ? 37 : (pos == 37 ? 699 : 700)) {
        for (u32 i = lane; i < 832; i += 64) big[i] = i < 700 ? (u64)(5000 - 3 * i) << 32 : 0;
        wave_sync();
        shift_up(big, pos, 700);
        st_one(big, pos, (u64)12345);
        wave_sync();
        for (u32 i = 0; i < 701; i++) {
            u64 want = i < pos ? (u64)(5000 - 3 * i) << 32 : (i == pos ? (u64)12345 : (u64)(5000 - 3 * (i - 1)) << 32);
            if (big[i] != want) bad |= 1024;
        }
        for (u32 i = 701; i < 832; i++)
            if (big[i] != 0) bad |= 1024;
        shift_down(big, pos, 701);
        for (u32 i = 0; i < 700; i++)
            if (big[i] != (u64)(5000 - 3 * i) << 32) bad |= 2048;
        for (u32 i = 701; i < 832; i++)
            if (big[i] != 0) bad |= 2048;
    }
    // arrays of narrow keys: block moves and the rank search with 128 probes in registers
    for (u32 n = 5; n <= 1900; n = n < 40 ? n + 1 : n * 3 + 7) {
        for (u32 pos = 0; pos < n; pos = pos < 18 ? pos + 1 : pos * 2 + 3) {
            for (u32 i = lane; i < 2048; i += 64) nar[i] = nar32[i] = i < n ? 4000 - 2 * i : 0;
            wave_sync();
            blk_shift_up(nar, pos, n);
            blk_shift_up(nar32, pos, n);
            st_one(nar, pos, (uint16_t)7);
            st_one(nar32, pos, 7u);
            wave_sync();
            for (u32 i = lane; i < 2048; i += 64) {
                const u32 want = i < pos ? 4000 - 2 * i : (i == pos ? 7u : (i <= n ? 4000 - 2 * (i - 1) : 0u));
                if (nar[i] != want || nar32[i] != want) bad |= 4096;
            }
            wave_sync();
            blk_shift_down(nar, pos, n + 1);
            blk_shift_down(nar32, pos, n + 1);
            for (u32 i = lane; i < 2048; i += 64) {
                const u32 want = i < n ? 4000 - 2 * i : 0u;
                if (nar[i] != want || nar32[i] != want) bad |= 8192;
            }
            wave_sync();
        }
        Probe2<uint16_t> pr;
        pr.refresh(nar, n);
        for (u32 key = 150; key <= 4003; key += 7) {
            u32 ref = 0;
            for (u32 i = 0; i < n; i++) ref += nar[i] > key ? 1u : 0u;
            if (pr.rank(nar, (uint16_t)key) != ref || rank_desc_k(nar, n, (uint16_t)key) != ref ||
                rank_desc_k(nar32, n, key) != ref)
                bad |= 16384;
            const u32 b0 = pr.block((uint16_t)key);
            if (b0 > ref || ref - b0 >= 64) bad |= 32768;
        }
    }
    u64 any = ballot(bad != 0);
    if (lane == 0) *fail = any ? (bad | 0x80000000u) : 0;
    if (any && bad) atomicOr(fail, bad);
}
