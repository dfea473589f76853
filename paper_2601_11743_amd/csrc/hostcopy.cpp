// Host-side byte movers: streaming copy for the pageable leg and the 64-bit hash.
//
// Paper, "Speeding Up Context Switches": the pageable<->pinned leg is copied by several
// threads so that DRAM bandwidth, not one core, is the limit.  Each copy here streams past the
// cache with non-temporal stores: the data is touched once and the destination line is never
// read first.
#include <immintrin.h>

#include <algorithm>
#include <atomic>
#include <cstring>
#include <thread>

#include "internal.hpp"

namespace nixie {

namespace {

__attribute__((target("avx2"))) void copy_stream_avx2(uint8_t *d, const uint8_t *s, size_t n) {
    size_t head = (32 - ((uintptr_t)d & 31)) & 31;
    if (head > n) head = n;
    if (head) { std::memcpy(d, s, head); d += head; s += head; n -= head; }
    size_t blocks = n / 128;
    for (size_t i = 0; i < blocks; i++) {
        __m256i a = _mm256_loadu_si256((const __m256i *)(s));
        __m256i b = _mm256_loadu_si256((const __m256i *)(s + 32));
        __m256i c = _mm256_loadu_si256((const __m256i *)(s + 64));
        __m256i e = _mm256_loadu_si256((const __m256i *)(s + 96));
        _mm256_stream_si256((__m256i *)(d), a);
        _mm256_stream_si256((__m256i *)(d + 32), b);
        _mm256_stream_si256((__m256i *)(d + 64), c);
        _mm256_stream_si256((__m256i *)(d + 96), e);
        s += 128;
        d += 128;
    }
    n -= blocks * 128;
    if (n) std::memcpy(d, s, n);
}

const bool g_have_avx2 = __builtin_cpu_supports("avx2");

}  // namespace

// The caller issues one store fence after the last copy of a batch (the stores here are
// weakly ordered).
void copy_stream(void *dst, const void *src, size_t n) {
    if (n < 512 || !g_have_avx2) {
        std::memcpy(dst, src, n);
        return;
    }
    copy_stream_avx2((uint8_t *)dst, (const uint8_t *)src, n);
}

uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Sum of the word terms k in [word_begin, word_end) of a buffer of n bytes (no length term).
uint64_t hash_host_range(const uint8_t *base, uint64_t n, uint64_t word_begin, uint64_t word_end) {
    constexpr uint64_t G = 0x9E3779B97F4A7C15ull;
    uint64_t acc = 0;
    uint64_t full = n / 8;
    uint64_t k = word_begin;
    for (; k < word_end && k < full; k++) {
        uint64_t w;
        std::memcpy(&w, base + 8 * k, 8);
        acc += mix64(w + G * (k + 1));
    }
    if (k < word_end) {  // the zero-padded last word
        uint64_t w = 0;
        std::memcpy(&w, base + 8 * k, (size_t)(n - 8 * k));
        acc += mix64(w + G * (k + 1));
    }
    return acc;
}

int hash_host_buffers(const void *const *ptrs, const uint64_t *bytes, uint64_t n, uint64_t *hashes,
                      unsigned threads) {
    constexpr uint64_t kUnitWords = 1u << 17;  // 1 MiB of input per work unit
    std::vector<uint64_t> first(n + 1, 0);
    for (uint64_t i = 0; i < n; i++) {
        if (bytes[i] && !ptrs[i]) return NIXIE_EINVAL;
        uint64_t words = (bytes[i] + 7) / 8;
        first[i + 1] = first[i] + (words + kUnitWords - 1) / kUnitWords;
        hashes[i] = mix64(bytes[i]);
    }
    const uint64_t units = first[n];
    if (units == 0) return NIXIE_OK;
    std::vector<std::atomic<uint64_t>> acc(n);
    for (auto &a : acc) a.store(0, std::memory_order_relaxed);
    std::atomic<uint64_t> next{0};
    auto work = [&]() {
        for (;;) {
            uint64_t u = next.fetch_add(1, std::memory_order_relaxed);
            if (u >= units) break;
            uint64_t i = (uint64_t)(std::upper_bound(first.begin(), first.end(), u) - first.begin()) - 1;
            uint64_t words = (bytes[i] + 7) / 8;
            uint64_t wb = (u - first[i]) * kUnitWords, we = std::min(words, wb + kUnitWords);
            acc[i].fetch_add(hash_host_range((const uint8_t *)ptrs[i], bytes[i], wb, we), std::memory_order_relaxed);
        }
    };
    unsigned T = (unsigned)std::min<uint64_t>(std::max(1u, threads), units);
    std::vector<std::thread> pool;
    for (unsigned t = 1; t < T; t++) pool.emplace_back(work);
    work();
    for (auto &t : pool) t.join();
    for (uint64_t i = 0; i < n; i++) hashes[i] += acc[i].load(std::memory_order_relaxed);
    return NIXIE_OK;
}

// dst[i][0..bytes[i]) = src[i][0..bytes[i]) for every i, in 1 MiB units handed to `threads` threads.
int copy_host_buffers(void *const *dst, const void *const *src, const uint64_t *bytes, uint64_t n, unsigned threads) {
    constexpr uint64_t kUnit = 1u << 20;
    std::vector<uint64_t> first(n + 1, 0);
    for (uint64_t i = 0; i < n; i++) {
        if (bytes[i] && (!dst[i] || !src[i])) return NIXIE_EINVAL;
        first[i + 1] = first[i] + (bytes[i] + kUnit - 1) / kUnit;
    }
    const uint64_t units = first[n];
    if (units == 0) return NIXIE_OK;
    std::atomic<uint64_t> next{0};
    auto work = [&]() {
        for (;;) {
            const uint64_t u = next.fetch_add(1, std::memory_order_relaxed);
            if (u >= units) break;
            const uint64_t i = (uint64_t)(std::upper_bound(first.begin(), first.end(), u) - first.begin()) - 1;
            const uint64_t b = (u - first[i]) * kUnit, e = std::min(bytes[i], b + kUnit);
            copy_stream((uint8_t *)dst[i] + b, (const uint8_t *)src[i] + b, e - b);
        }
        _mm_sfence();
    };
    const unsigned T = (unsigned)std::min<uint64_t>(std::max(1u, threads), units);
    std::vector<std::thread> pool;
    for (unsigned t = 1; t < T; t++) pool.emplace_back(work);
    work();
    for (auto &t : pool) t.join();
    return NIXIE_OK;
}

}  // namespace nixie
