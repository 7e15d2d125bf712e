// Dense row gather: out row i <- the bytes of a source row chosen per i.
//
// The output is treated as one flat, dense stream, whatever the row length.
// Two kernels:
//   * gather_chunks_kernel (rows a multiple of 4 bytes, 16-byte aligned
//     output): every thread produces 16 consecutive output bytes with one
//     aligned 16-byte non-temporal store. The 16 bytes normally come from one
//     source row and are read with a single 16-byte load that only needs 4-byte
//     alignment; a thread whose bytes straddle a row end falls back to 4-byte
//     loads. A wave instruction therefore moves 1 KiB, rows of any length
//     (372 B, 1652 B, ...) fill every lane, and the dense output is written in
//     whole 128-byte lines.
//   * gather_elems_kernel: the same flat scheme with one V-wide element (2, 4,
//     8 or 16 bytes) per thread, for rows or bases that are only 2-byte aligned.
// Where a row comes from is a functor, so the kernels serve both a table in
// device memory and the cache's choice of cache row / staged row / host row.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace taser_gather {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <typename V> __device__ __forceinline__ V zero_of() { return V(0); }
template <> __device__ __forceinline__ u32x4 zero_of<u32x4>() { return u32x4{0, 0, 0, 0}; }
template <> __device__ __forceinline__ u32x2 zero_of<u32x2>() { return u32x2{0, 0}; }

constexpr int kThreads = 256;
constexpr int kUnroll = 4;
constexpr int kTile = kThreads * kUnroll;   // elements (or 16-byte chunks) per block
constexpr int kMaxTileRows = kTile * 4 + 2; // output rows a block of the chunk kernel can touch (rows of one dword)

// 16 bytes that are only known to be 4-byte aligned.
struct __attribute__((packed, aligned(4))) Chunk16 {
    u32x4 v;
};

typedef const __attribute__((address_space(1))) Chunk16* GlobalChunk16Ptr;
typedef const __attribute__((address_space(1))) uint32_t* GlobalU32Ptr;

// A Source says where output row i comes from, in two steps so that the kernel
// can issue the (dependent) loads of several rows back to back:
//   key(i)          a 32-bit token read from memory (an id, a cache location);
//   address(key, i) first byte of the source row, or nullptr for a zero row.
// row(i) is the two combined.

// USE_MAGIC: floor(e / d) = umulhi(e, magic) with magic = ceil(2^32 / d), exact
// for e * d < 2^32 (the launcher checks that); otherwise a plain division.
template <typename Source, bool USE_MAGIC>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void gather_chunks_kernel(Source source, uint32_t row_dwords, uint32_t magic,
                                                                 int64_t total_dwords, int64_t last_row,
                                                                 const uint8_t* __restrict__ zeros,
                                                                 uint32_t* __restrict__ out) {
    const int64_t tile = (int64_t)blockIdx.x * (kTile * 4);   // first output dword of this block
    int64_t row0;                                               // output row holding it
    if (tile < ((int64_t)1 << 32)) row0 = (uint32_t)tile / row_dwords;
    else row0 = tile / (int64_t)row_dwords;
    const uint32_t col0 = (uint32_t)(tile - row0 * row_dwords);

    // Pass 0: the tokens of every output row this tile touches, loaded once by consecutive
    // lanes into LDS. Without it each chunk's token is a wave-wide broadcast load at the head of
    // a chain of two dependent loads, and the kernel's speed follows the latency of the token
    // array (slower by a third when that array has dropped out of the memory-side cache).
    __shared__ int32_t tile_key[kMaxTileRows];
    {
        int64_t tile_last = tile + kTile * 4 - 1;
        if (tile_last >= total_dwords) tile_last = total_dwords - 1;
        const uint32_t e_last = col0 + (uint32_t)(tile_last - tile);   // dword offset from the start of row0
        const int rows_here = (int)(USE_MAGIC ? __umulhi(e_last, magic) : e_last / row_dwords) + 1;   // <= kMaxTileRows
        for (int r = threadIdx.x; r < rows_here; r += kThreads) tile_key[r] = source.key(row0 + r);
        __syncthreads();
    }
    // Pass 1 (ALU only): output row and column of each of this thread's chunks.
    uint32_t col[kUnroll];
    int64_t row[kUnroll];
    bool whole[kUnroll], cross[kUnroll];   // inside one row / crossing a row end (neither: past the end)
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint32_t local = (threadIdx.x + u * kThreads) * 4u;
        const uint32_t e = col0 + local;                        // dword offset from the start of row0
        const uint32_t dr = USE_MAGIC ? __umulhi(e, magic) : e / row_dwords;
        col[u] = e - dr * row_dwords;
        row[u] = row0 + dr;
        const bool live = tile + local < total_dwords;
        whole[u] = live && col[u] + 4u <= row_dwords;
        cross[u] = live && !whole[u];
        if (row[u] > last_row) row[u] = last_row;               // keeps the token read below in bounds
    }
    // Pass 2: straight-line code, no branches, so that the four 16-byte row loads are in
    // flight together. A chunk with nothing to load here (zero row, row-crossing, past the
    // end) reads 16 zero bytes instead of branching around the load.
    int32_t key[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) key[u] = tile_key[row[u] - row0];
    u32x4 vals[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint8_t* base = source.address(key[u], row[u]);
        const uint8_t* at = (whole[u] && base) ? base + (size_t)col[u] * 4u : zeros;
        vals[u] = ((GlobalChunk16Ptr)at)->v;
    }
    // Pass 3 (rare): chunks that cross one or more row ends, dword by dword.
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        if (!cross[u]) continue;
        const int64_t d = tile + (threadIdx.x + u * kThreads) * 4u;
        uint32_t c = col[u];
        int64_t r = row[u];
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (c >= row_dwords) { c = 0; ++r; }
            if (d + i < total_dwords) {
                const uint8_t* base = source.address(tile_key[r - row0], r);
                if (base) w[i] = ((GlobalU32Ptr)base)[c];
            }
            ++c;
        }
        vals[u] = u32x4{w[0], w[1], w[2], w[3]};
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t d = tile + (threadIdx.x + u * kThreads) * 4u;
        if (d + 4 <= total_dwords) {
            __builtin_nontemporal_store(vals[u], reinterpret_cast<u32x4*>(out + d));
        } else {
            const uint32_t w[4] = {vals[u].x, vals[u].y, vals[u].z, vals[u].w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (d + i < total_dwords) out[d + i] = w[i];
        }
    }
}

// ---- gather with source rows owned by L2 partitions ------------------------------
// The chip's L2 is split over kOwnerClasses dies, each caching what its own compute
// units read; workgroups go to the dies round-robin, so workgroup b runs on die
// b % kOwnerClasses. A source table a few times larger than one die's L2 but smaller
// than all of them together is re-read from memory again and again when every
// workgroup may read every row. Here a Source also gives every request an owner class,
// a function of the source row (so that one die reads a row, and only it), or of the
// request's position for rows so popular that they sit in every L2 anyway.
// Work is handed out in output lines of 128 bytes: a line belongs to the class of the
// output row that holds its first byte, so every line is written whole by one workgroup.
// kOwnerClasses workgroups look at the same super-tile of kOwnedTileLines lines; each
// lists the rows of its class (all per-row arithmetic done once per row, into LDS) and
// spreads the 16-byte chunks of their lines over its lanes. The chunks of a row's last
// line that lie beyond the row's end belong to the next output row and are read there.
// The assumption about where workgroups run only affects speed, never results.
constexpr int kOwnerClasses = 8;
constexpr int kOwnedTileLines = 1536;     // 192 KiB of output per super-tile: about 1500 chunks per workgroup; smaller
                                          // tiles leave the workgroups' shares too uneven, larger ones cost LDS
constexpr int kOwnedMinRowBytes = 512;
constexpr int kOwnedMaxRowBytes = 16384;
constexpr int kOwnedMaxRows = kOwnedTileLines * 128 / kOwnedMinRowBytes + 3;

template <typename Source>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void gather_owned_lines_kernel(
    Source source, uint32_t row_bytes, uint32_t slots, uint32_t slot_magic, uint32_t step_rows, uint32_t step_rest,
    int64_t total_bytes, int64_t n_rows, const uint8_t* __restrict__ zeros, uint8_t* __restrict__ out) {
    __shared__ int32_t tile_key[kOwnedMaxRows + 1];
    __shared__ const uint8_t* own_base[kOwnedMaxRows];   // source row, or `zeros` with the zero flag set
    __shared__ const uint8_t* own_next[kOwnedMaxRows];   // source row of the next output row minus row_bytes (same flag rule)
    __shared__ uint32_t own_meta[kOwnedMaxRows];          // first line in the tile + 256 | lines << 12 | bytes before the first line << 20
                                                          // | bit 30: this row is zeros | bit 31: the next row is zeros
    __shared__ uint32_t n_owned;

    const uint32_t cls = blockIdx.x % kOwnerClasses;
    const int64_t line0 = (int64_t)(blockIdx.x / kOwnerClasses) * kOwnedTileLines;
    const int64_t total_lines = (total_bytes + 127) >> 7;
    const uint32_t lines_here = (uint32_t)(total_lines - line0 < kOwnedTileLines ? total_lines - line0 : kOwnedTileLines);
    const int64_t tile_byte0 = line0 * 128;
    const uint32_t tile_limit = (uint32_t)(total_bytes - tile_byte0 < (int64_t)kOwnedTileLines * 128 ? total_bytes - tile_byte0
                                                                                                  : (int64_t)kOwnedTileLines * 128);
    const int64_t r0 = tile_byte0 / row_bytes;                              // row holding the tile's first byte
    int64_t r_last = (tile_byte0 + (int64_t)lines_here * 128 - 1) / row_bytes;   // row holding its last byte
    if (r_last > n_rows - 1) r_last = n_rows - 1;
    const int rows_here = (int)(r_last - r0 + 1);                           // <= kOwnedMaxRows - 1
    const int keys_here = rows_here + (r_last + 1 < n_rows ? 1 : 0);        // + the row the last line may run into
    if (threadIdx.x == 0) n_owned = 0;
    for (int i = threadIdx.x; i < keys_here; i += kThreads) tile_key[i] = source.key(r0 + i);
    __syncthreads();
    for (int i = threadIdx.x; i < rows_here; i += kThreads) {
        const int64_t r = r0 + i;
        const int32_t key = tile_key[i];
        if (source.owner(key, r) != cls) continue;
        const int64_t begin = r * row_bytes;
        const int64_t first = (begin + 127) >> 7, next = (begin + row_bytes + 127) >> 7;   // lines whose first byte is in row r
        const uint8_t* base = source.address(key, r);
        const uint8_t* after = i + 1 < keys_here ? source.address(tile_key[i + 1], r + 1) : nullptr;
        const uint32_t at = atomicAdd(&n_owned, 1u);
        own_base[at] = base ? base : zeros;
        own_next[at] = after ? after - row_bytes : zeros;
        own_meta[at] = (uint32_t)(first - line0 + 256) | ((uint32_t)(next - first) << 12) | ((uint32_t)(first * 128 - begin) << 20) |
                       (base ? 0u : 1u << 30) | (after ? 0u : 1u << 31);
    }
    __syncthreads();

    const uint32_t items = n_owned * slots;          // `slots` 16-byte chunks per owned row, some of them beyond its lines
    for (uint32_t round = 0; round < items; round += kTile) {
        const uint8_t* from[kUnroll];
        uint32_t out_off[kUnroll], which[kUnroll], in_off[kUnroll];
        bool whole[kUnroll], cross[kUnroll];
        // one division per thread: its further chunks lie kThreads = step_rows * slots + step_rest chunks on
        const uint32_t w0 = round + threadIdx.x;
        uint32_t j = __umulhi(w0, slot_magic), within = w0 - j * slots;   // exact: w0 * slots < 2^32
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const bool live = round + threadIdx.x + u * kThreads < items;
            const uint32_t jj = live ? j : 0u;
            const uint32_t meta = own_meta[jj];
            const uint32_t line = (meta & 4095u) + (within >> 3) - 256u;          // relative to the tile; wraps if before it
            const bool mine = live && (within >> 3) < ((meta >> 12) & 255u) && line < lines_here;
            out_off[u] = line * 128u + (within & 7u) * 16u;
            uint32_t off = ((meta >> 20) & 255u) + within * 16u;                   // bytes from the row's start
            const bool beyond = off >= row_bytes;                                  // the chunk lies in the next output row
            const uint8_t* base = beyond ? own_next[jj] : own_base[jj];
            const bool zero = (meta >> (beyond ? 31 : 30)) & 1u;
            whole[u] = mine && out_off[u] + 16u <= tile_limit && (beyond || off + 16u <= row_bytes);
            cross[u] = mine && !whole[u] && out_off[u] < tile_limit;
            from[u] = (whole[u] && !zero) ? base + off : zeros;
            in_off[u] = off;
            which[u] = jj;
            j += step_rows;
            within += step_rest;
            if (within >= slots) {
                within -= slots;
                ++j;
            }
        }
        u32x4 vals[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) vals[u] = ((GlobalChunk16Ptr)from[u])->v;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (!cross[u]) continue;
            // dword by dword: the rest of the row, then the start of the next one (or the output's ragged end)
            const uint32_t meta = own_meta[which[u]];
            const uint8_t *a = own_base[which[u]], *b = own_next[which[u]];
            uint32_t wds[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t off = in_off[u] + 4u * e;
                if (out_off[u] + 4u * e >= tile_limit) continue;
                const bool beyond = off >= row_bytes;
                const bool zero = (meta >> (beyond ? 31 : 30)) & 1u;
                if (!zero) wds[e] = *(GlobalU32Ptr)((beyond ? b : a) + off);
            }
            vals[u] = u32x4{wds[0], wds[1], wds[2], wds[3]};
        }
        uint8_t* tile_out = out + tile_byte0;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            if (whole[u] || (cross[u] && out_off[u] + 16u <= tile_limit)) {
                __builtin_nontemporal_store(vals[u], reinterpret_cast<u32x4*>(tile_out + out_off[u]));
            } else if (cross[u]) {
                const uint32_t wds[4] = {vals[u].x, vals[u].y, vals[u].z, vals[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (out_off[u] + 4u * e < tile_limit) reinterpret_cast<uint32_t*>(tile_out + out_off[u])[e] = wds[e];
            }
        }
    }
}

template <typename V, typename Source>
__global__ __launch_bounds__(kThreads) void gather_elems_kernel(Source source, uint32_t row_elems,
                                                                int64_t total_elems, V* __restrict__ out) {
    const int64_t tile = (int64_t)blockIdx.x * kTile;
    int64_t row0;
    if (tile < ((int64_t)1 << 32)) row0 = (uint32_t)tile / row_elems;
    else row0 = tile / (int64_t)row_elems;
    const uint32_t col0 = (uint32_t)(tile - row0 * row_elems);

    V vals[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const uint32_t e = col0 + threadIdx.x + u * kThreads;
        const uint32_t dr = e / row_elems;
        const uint32_t col = e - dr * row_elems;
        const int64_t g = tile + threadIdx.x + u * kThreads;
        vals[u] = zero_of<V>();
        if (g < total_elems) {
            const int64_t row = row0 + dr;
            const uint8_t* base = source.address(source.key(row), row);
            if (base) vals[u] = reinterpret_cast<const V*>(base)[col];
        }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
        const int64_t g = tile + threadIdx.x + u * kThreads;
        if (g < total_elems) __builtin_nontemporal_store(vals[u], out + g);
    }
}

// Largest power-of-two width (16, 8, 4, 2 or 1) dividing everything given.
inline int common_alignment(uint64_t bits) {
    if ((bits & 15) == 0) return 16;
    if ((bits & 7) == 0) return 8;
    if ((bits & 3) == 0) return 4;
    if ((bits & 1) == 0) return 2;
    return 1;
}

template <typename V, typename Source>
inline void launch_elems(const Source& source, int32_t row_bytes, int64_t n, void* out, hipStream_t stream) {
    const uint32_t row_elems = (uint32_t)(row_bytes / (int)sizeof(V));
    const int64_t total = n * (int64_t)row_elems;
    const int64_t blocks = (total + kTile - 1) / kTile;
    hipLaunchKernelGGL((gather_elems_kernel<V, Source>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, source,
                       row_elems, total, reinterpret_cast<V*>(out));
}

// Device address of 16 zero bytes (defined once, in gather.hip); nullptr on failure.
const uint8_t* zero_chunk();

// `src_align`: power of two dividing the row size, every source pitch and every
// source base address. Returns false if the launch would need more blocks than
// a grid dimension holds.
template <typename Source>
inline bool launch(const Source& source, int src_align, int32_t row_bytes, int64_t n, void* out, hipStream_t stream) {
    if (n == 0) return true;
    const uint8_t* zeros = zero_chunk();
    if (!zeros) return false;
    const uint64_t out_bits = (uint64_t)(uintptr_t)out;
    if (src_align >= 4 && (out_bits & 15) == 0) {
        const uint32_t row_dwords = (uint32_t)row_bytes / 4u;
        const int64_t total = n * (int64_t)row_dwords;
        const int64_t blocks = (total + kTile * 4 - 1) / (kTile * 4);
        if (blocks > 0x7fffffffLL) return false;
        // the in-block offsets stay below row_dwords + 4 * kTile: exact while that is < 2^32 / row_dwords
        const bool small = (uint64_t)row_dwords * ((uint64_t)row_dwords + 4u * kTile) < ((uint64_t)1 << 32);
        if (small && row_dwords > 1) {
            const uint32_t magic = (uint32_t)((((uint64_t)1 << 32) + row_dwords - 1) / row_dwords);
            hipLaunchKernelGGL((gather_chunks_kernel<Source, true>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                               source, row_dwords, magic, total, n - 1, zeros, reinterpret_cast<uint32_t*>(out));
        } else {
            hipLaunchKernelGGL((gather_chunks_kernel<Source, false>), dim3((unsigned)blocks), dim3(kThreads), 0, stream,
                               source, row_dwords, 0u, total, n - 1, zeros, reinterpret_cast<uint32_t*>(out));
        }
        return true;
    }
    const int align = common_alignment((uint64_t)src_align | out_bits);
    const int64_t total = n * (int64_t)(row_bytes / align);
    if ((total + kTile - 1) / kTile > 0x7fffffffLL) return false;
    switch (align) {
        case 16: launch_elems<u32x4>(source, row_bytes, n, out, stream); break;
        case 8: launch_elems<u32x2>(source, row_bytes, n, out, stream); break;
        case 4: launch_elems<uint32_t>(source, row_bytes, n, out, stream); break;
        default: launch_elems<uint16_t>(source, row_bytes, n, out, stream); break;
    }
    return true;
}

// The same for a Source that also has owner(key, i) (see gather_owned_lines_kernel), used when
// the rows are long enough and the request count large enough for it to pay; otherwise, and for
// an output that is not 16-byte aligned, this is launch().
template <typename Source>
inline bool launch_owned(const Source& source, int src_align, int32_t row_bytes, int64_t n, void* out, hipStream_t stream) {
    const uint64_t out_bits = (uint64_t)(uintptr_t)out;
    if (src_align < 4 || (out_bits & 15) || row_bytes < kOwnedMinRowBytes || row_bytes > kOwnedMaxRowBytes || n < 4096)
        return launch(source, src_align, row_bytes, n, out, stream);
    const uint8_t* zeros = zero_chunk();
    if (!zeros) return false;
    const int64_t total_bytes = n * (int64_t)row_bytes;
    const uint32_t slots = (uint32_t)((row_bytes + 127) / 128) * 8u;       // chunks of the most lines a row can own
    // items of a workgroup stay far below 2^32 / slots: the multiply-high division is exact
    const uint32_t slot_magic = (uint32_t)((((uint64_t)1 << 32) + slots - 1) / slots);
    const int64_t tiles = ((total_bytes + 127) / 128 + kOwnedTileLines - 1) / kOwnedTileLines;
    if (tiles * kOwnerClasses > 0x7fffffffLL) return false;
    hipLaunchKernelGGL((gather_owned_lines_kernel<Source>), dim3((unsigned)(tiles * kOwnerClasses)), dim3(kThreads), 0, stream,
                       source, (uint32_t)row_bytes, slots, slot_magic, (uint32_t)kThreads / slots, (uint32_t)kThreads % slots,
                       total_bytes, n, zeros, static_cast<uint8_t*>(out));
    return true;
}

}  // namespace taser_gather
