/*
 * randline_oracle.c -- CPU oracle for the random cache-line read benchmark.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and the
 * product never calls it; only the tests, the smoke check and the CPU-baseline
 * leg of the benchmark driver load it.
 *
 * What the benchmark is (paper, Sec. 1.3 and Sec. 2.1): every warp repeatedly
 * picks a random, aligned, coalesced line (32 words of 32 bits = 128 bytes;
 * Sec. 2.1 also quotes 32 x 64-bit and 32 x 128-bit lines) anywhere in a memory
 * region of a chosen size and reads it.  Optionally (Sec. 2.1 second experiment,
 * Sec. 2.4) the region is cut into equal chunks and all warps of one compute
 * group read only from that group's chunk.
 *
 * The paper measures time only.  To make "the right lines were read" checkable
 * the build adds a checksum, and that is what this oracle computes:
 *
 *   - the region holds a known pseudo-random fill (fill_word below);
 *   - logical wave w, iteration it, reads the line with index
 *         window_base(w) + H(read_seed, w, it) mod L_win ;
 *   - the checksum is the sum modulo 2^64 of every 32-bit word (zero extended)
 *     of every line read.
 *
 * The paper fixes none of the generator details; the readings taken here are:
 *   mix64      : output function of the SplitMix64 generator (Steele, Lea,
 *                Flood, "Fast splittable pseudorandom number generators", 2014).
 *   sm(s,k)    : k-th output (k = 0,1,..) of SplitMix64 seeded with s,
 *                i.e. mix64(s + (k+1)*GAMMA).
 *   fill       : the region viewed as little-endian uint64[R/8] is the SplitMix64
 *                stream of fill_seed: u64[j] = sm(fill_seed, j).  32-bit word i is
 *                the low (i even) or high (i odd) half of u64[i/2].
 *   H(s,w,it)  : sm(sm(s,w), it) -- one generator per logical wave, split off
 *                the read seed; iteration it takes its it-th output.
 *   reduction  : exact unsigned remainder modulo the number of lines in the window.
 *   windows    : n_windows equal, disjoint, contiguous chunks of L/n_windows lines;
 *                logical wave w belongs to group w mod G and reads only from
 *                chunk window_of_group[w mod G].
 *
 * Two independent evaluation modes are provided so that each checks the other:
 *   recompute    : never touches a buffer, regenerates each word from its index;
 *   materialised : fills a real host buffer and performs the reads from memory.
 *
 * All arithmetic is on uint64_t / uint32_t and wraps.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define RLO_OK 0
#define RLO_EINVAL (-1)

static const uint64_t GAMMA = 0x9E3779B97F4A7C15ULL; /* SplitMix64 increment */

/* SplitMix64 output function. */
uint64_t rlo_mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* k-th output (0-based) of a SplitMix64 generator whose state starts at s. */
uint64_t rlo_sm(uint64_t s, uint64_t k) {
    return rlo_mix64(s + (k + 1) * GAMMA);
}

/* Content of 32-bit word number i of a region filled with fill_seed. */
uint32_t rlo_fill_word(uint64_t fill_seed, uint64_t i) {
    uint64_t q = rlo_sm(fill_seed, i / 2);
    return (i % 2 == 0) ? (uint32_t)(q & 0xFFFFFFFFULL) : (uint32_t)(q >> 32);
}

/* Raw 64-bit draw of logical wave w at iteration it. */
uint64_t rlo_index_hash(uint64_t read_seed, uint64_t w, uint64_t it) {
    uint64_t wave_seed = rlo_sm(read_seed, w);
    return rlo_sm(wave_seed, it);
}

/* Argument checks shared by the entry points below. */
static int check_args(uint64_t region_bytes, uint32_t line_bytes, uint32_t G,
                      uint32_t n_windows, const uint16_t *window_of_group) {
    if (line_bytes != 128 && line_bytes != 256 && line_bytes != 512) return RLO_EINVAL;
    if (region_bytes == 0 || region_bytes % line_bytes != 0) return RLO_EINVAL;
    if (G == 0 || n_windows == 0) return RLO_EINVAL;
    uint64_t L = region_bytes / line_bytes;
    if (L % n_windows != 0) return RLO_EINVAL;
    if (G > 1 || n_windows > 1) {
        if (window_of_group == NULL) return RLO_EINVAL;
        for (uint32_t g = 0; g < G; ++g)
            if (window_of_group[g] >= n_windows) return RLO_EINVAL;
    }
    return RLO_OK;
}

/* Line index (within the whole region) read by logical wave w at iteration it. */
static uint64_t line_of(uint64_t read_seed, uint64_t w, uint64_t it, uint64_t L,
                        uint32_t G, uint32_t n_windows, const uint16_t *window_of_group) {
    uint64_t L_win = L / n_windows;
    uint64_t window = (window_of_group != NULL) ? window_of_group[w % G] : 0;
    return window * L_win + rlo_index_hash(read_seed, w, it) % L_win;
}

/*
 * Write the line indices of logical waves [first_wave, first_wave+W), I
 * iterations each, into out[(w-first_wave)*I + it].  For tests of range and
 * uniformity.
 */
int rlo_indices(uint64_t region_bytes, uint32_t line_bytes, uint64_t first_wave, uint64_t W,
                uint32_t I, uint32_t G, uint32_t n_windows, const uint16_t *window_of_group,
                uint64_t read_seed, uint64_t *out) {
    int rc = check_args(region_bytes, line_bytes, G, n_windows, window_of_group);
    if (rc != RLO_OK || out == NULL) return RLO_EINVAL;
    uint64_t L = region_bytes / line_bytes;
    for (uint64_t a = 0; a < W; ++a)
        for (uint64_t it = 0; it < I; ++it)
            out[a * I + it] = line_of(read_seed, first_wave + a, it, L, G, n_windows, window_of_group);
    return RLO_OK;
}

/*
 * Recompute mode.  Checksum of logical waves [first_wave, first_wave+W), I
 * iterations each.  n_threads <= 1 runs serially; otherwise the wave range is
 * split over that many threads (the sum is commutative, so the split cannot
 * change the value).  *threads_used reports how many threads actually ran.
 */
int rlo_checksum(uint64_t region_bytes, uint32_t line_bytes, uint64_t first_wave, uint64_t W,
                 uint32_t I, uint32_t G, uint32_t n_windows, const uint16_t *window_of_group,
                 uint64_t fill_seed, uint64_t read_seed, int n_threads, uint64_t *checksum,
                 int *threads_used) {
    int rc = check_args(region_bytes, line_bytes, G, n_windows, window_of_group);
    if (rc != RLO_OK || checksum == NULL) return RLO_EINVAL;
    uint64_t L = region_bytes / line_bytes;
    uint64_t words_per_line = line_bytes / 4;
    uint64_t total = 0;
    int used = 1;
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) reduction(+ : total) schedule(static)
#endif
    for (int64_t a = 0; a < (int64_t)W; ++a) {
#ifdef _OPENMP
        if (a == 0) used = omp_get_num_threads();
#endif
        uint64_t w = first_wave + (uint64_t)a;
        uint64_t wave_sum = 0;
        for (uint64_t it = 0; it < I; ++it) {
            uint64_t line = line_of(read_seed, w, it, L, G, n_windows, window_of_group);
            uint64_t first_word = line * words_per_line;
            for (uint64_t j = 0; j < words_per_line; ++j)
                wave_sum += (uint64_t)rlo_fill_word(fill_seed, first_word + j);
        }
        total += wave_sum;
    }
    *checksum = total;
    if (threads_used) *threads_used = used;
    return RLO_OK;
}

/* Materialise the fill into a host buffer of `bytes` bytes (multiple of 8). */
int rlo_fill_buffer(void *buf, uint64_t bytes, uint64_t fill_seed) {
    if (buf == NULL || bytes % 8 != 0) return RLO_EINVAL;
    unsigned char *p = (unsigned char *)buf;
    for (uint64_t j = 0; j < bytes / 8; ++j) {
        uint64_t q = rlo_sm(fill_seed, j);
        for (int b = 0; b < 8; ++b) p[8 * j + b] = (unsigned char)(q >> (8 * b)); /* little endian */
    }
    return RLO_OK;
}

/*
 * Materialised mode.  Same checksum, but every word is actually loaded from
 * `buf` (region_bytes long, any content): this is the host-memory analogue of
 * the benchmark, and with a buffer produced by rlo_fill_buffer it must agree
 * with rlo_checksum.
 */
int rlo_checksum_materialised(const void *buf, uint64_t region_bytes, uint32_t line_bytes,
                              uint64_t first_wave, uint64_t W, uint32_t I, uint32_t G,
                              uint32_t n_windows, const uint16_t *window_of_group,
                              uint64_t read_seed, int n_threads, uint64_t *checksum,
                              int *threads_used) {
    int rc = check_args(region_bytes, line_bytes, G, n_windows, window_of_group);
    if (rc != RLO_OK || checksum == NULL || buf == NULL) return RLO_EINVAL;
    uint64_t L = region_bytes / line_bytes;
    const unsigned char *base = (const unsigned char *)buf;
    uint64_t total = 0;
    int used = 1;
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) reduction(+ : total) schedule(static)
#endif
    for (int64_t a = 0; a < (int64_t)W; ++a) {
#ifdef _OPENMP
        if (a == 0) used = omp_get_num_threads();
#endif
        uint64_t w = first_wave + (uint64_t)a;
        uint64_t wave_sum = 0;
        for (uint64_t it = 0; it < I; ++it) {
            uint64_t line = line_of(read_seed, w, it, L, G, n_windows, window_of_group);
            const unsigned char *p = base + line * (uint64_t)line_bytes;
            for (uint32_t off = 0; off < line_bytes; off += 4) {
                uint32_t word;
                memcpy(&word, p + off, 4); /* host is little endian, as is the GPU */
                wave_sum += (uint64_t)word;
            }
        }
        total += wave_sum;
    }
    *checksum = total;
    if (threads_used) *threads_used = used;
    return RLO_OK;
}

/* Fill words [first_word, first_word+n) into out[] -- for checking a GPU fill. */
int rlo_fill_words(uint64_t fill_seed, uint64_t first_word, uint64_t n, uint32_t *out) {
    if (out == NULL) return RLO_EINVAL;
    for (uint64_t k = 0; k < n; ++k) out[k] = rlo_fill_word(fill_seed, first_word + k);
    return RLO_OK;
}

/*
 * Streaming read: wrapping 64-bit sum of the 32-bit words [first_word,
 * first_word+n_words) of a region filled with fill_seed (zero extended).  The
 * definition of the sequential-read checksum; threads only split the range.
 */
int rlo_sum_words(uint64_t fill_seed, uint64_t first_word, uint64_t n_words, int n_threads,
                  uint64_t *sum) {
    if (sum == NULL) return RLO_EINVAL;
    uint64_t total = 0;
#ifdef _OPENMP
    if (n_threads < 1) n_threads = 1;
#pragma omp parallel for num_threads(n_threads) reduction(+ : total) schedule(static)
#endif
    for (int64_t k = 0; k < (int64_t)n_words; ++k)
        total += (uint64_t)rlo_fill_word(fill_seed, first_word + (uint64_t)k);
    *sum = total;
    return RLO_OK;
}

/*
 * Dependent-load walk (a latency probe in the spirit of the TLB-probing work
 * the paper cites in Sec. 1.3; the paper itself does not run one).  Starting at
 * line `start`, each hop loads 32-bit word 0 of the current line and moves to
 *     next = (line + stride + ((word ^ salt_k) & mask)) mod L ,   L = region_bytes/line_bytes,
 * where salt_k = (k * 0x9E3779B9) mod 2^32 for hop k = 0, 1, ...  The salt makes the step depend
 * on the hop number as well, so the walk is not the iteration of one fixed map and cannot fall
 * into a short cycle (which would sit in the caches).  mask = 0 gives a plain strided walk,
 * mask = 0xFFFFFFFF with stride 0 a data-driven pseudo-random walk.  Returns the line reached
 * after `hops` hops and the wrapping 64-bit sum of the words loaded on the way.
 */
int rlo_chase(uint64_t region_bytes, uint32_t line_bytes, uint64_t fill_seed, uint64_t start,
              uint64_t stride, uint32_t mask, uint64_t hops, uint64_t *final_line, uint64_t *word_sum) {
    if (line_bytes != 128 && line_bytes != 256 && line_bytes != 512) return RLO_EINVAL;
    if (region_bytes == 0 || region_bytes % line_bytes != 0) return RLO_EINVAL;
    if (final_line == NULL || word_sum == NULL) return RLO_EINVAL;
    uint64_t L = region_bytes / line_bytes;
    if (start >= L) return RLO_EINVAL;
    uint64_t words_per_line = line_bytes / 4;
    uint64_t line = start, sum = 0;
    for (uint64_t k = 0; k < hops; ++k) {
        uint32_t word = rlo_fill_word(fill_seed, line * words_per_line);
        sum += (uint64_t)word;
        uint32_t salt = (uint32_t)(k * 0x9E3779B9ULL);
        line = (line + stride % L + (uint64_t)((word ^ salt) & mask)) % L;
    }
    *final_line = line;
    *word_sum = sum;
    return RLO_OK;
}

/*
 * Random line write / read-modify-write (the other two access kinds of the
 * application the paper has in mind, Sec. 1.3; it measures reads only).  The
 * lines are those of the read benchmark without windows: logical wave w,
 * iteration it -> line H(draw_seed, w, it) mod L.  Every 32-bit word i of such a
 * line receives the value v(i) = low 32 bits of (value_seed + i * 0x9E3779B1):
 *   op 1 (write): word i = v(i);      op 2 (add): word i = word i + v(i) mod 2^32.
 * rlo_update_value      : v(i).
 * rlo_update_checksum   : wrapping 64-bit sum of v(i) over all words of all lines hit (repeats count).
 * rlo_apply_updates     : performs the updates, one after the other, on a host buffer.
 */
uint32_t rlo_update_value(uint64_t value_seed, uint64_t i) {
    return (uint32_t)((value_seed + i * 0x9E3779B1ULL) & 0xFFFFFFFFULL);
}

int rlo_update_checksum(uint64_t region_bytes, uint32_t line_bytes, uint64_t W, uint32_t I,
                        uint64_t draw_seed, uint64_t value_seed, uint64_t *checksum) {
    int rc = check_args(region_bytes, line_bytes, 1, 1, NULL);
    if (rc != RLO_OK || checksum == NULL) return RLO_EINVAL;
    uint64_t L = region_bytes / line_bytes, words_per_line = line_bytes / 4, total = 0;
    for (uint64_t w = 0; w < W; ++w)
        for (uint64_t it = 0; it < I; ++it) {
            uint64_t line = rlo_index_hash(draw_seed, w, it) % L;
            for (uint64_t j = 0; j < words_per_line; ++j)
                total += (uint64_t)rlo_update_value(value_seed, line * words_per_line + j);
        }
    *checksum = total;
    return RLO_OK;
}

int rlo_apply_updates(void *buf, uint64_t region_bytes, uint32_t line_bytes, uint64_t W, uint32_t I,
                      uint64_t draw_seed, uint32_t op, uint64_t value_seed) {
    int rc = check_args(region_bytes, line_bytes, 1, 1, NULL);
    if (rc != RLO_OK || buf == NULL || (op != 1 && op != 2)) return RLO_EINVAL;
    uint64_t L = region_bytes / line_bytes, words_per_line = line_bytes / 4;
    unsigned char *base = (unsigned char *)buf;
    for (uint64_t w = 0; w < W; ++w)
        for (uint64_t it = 0; it < I; ++it) {
            uint64_t line = rlo_index_hash(draw_seed, w, it) % L;
            for (uint64_t j = 0; j < words_per_line; ++j) {
                uint64_t i = line * words_per_line + j;
                uint32_t v = rlo_update_value(value_seed, i), old;
                memcpy(&old, base + 4 * i, 4);
                uint32_t now = (op == 1) ? v : (uint32_t)(old + v);
                memcpy(base + 4 * i, &now, 4);
            }
        }
    return RLO_OK;
}
