/*
 * bifeat_produce.hpp - fit and encode a table that is produced inside the kernels.
 *
 * bifeat_fit_update / bifeat_quantize read a chunk of the raw table from GPU memory.  When
 * the caller can make the values on the fly (a generator, a decoder of some other format, a
 * transformation of another array), the raw chunk need not exist at all: the two templates
 * below run the library's own fit and encode kernels over a caller-defined *row source*, so
 * that the one-time preprocessing (paper Sec. 3.3; Appendix D: one pass to fit, one to encode)
 * writes nothing but the packed codes.
 *
 * This is a C++/HIP interface: include it from a .hip file of your own, with the library's
 * csrc/ directory on the include path (the kernels are templates, instantiated in your
 * translation unit for your source type), and link against libbifeat.so for the bookkeeping
 * calls declared in bifeat.h (bifeat_produce_*).  Results are those of the chunk entry points
 * on a chunk holding the same values, bit for bit.
 *
 * A row source is any trivially copyable type with
 *     struct Ctx;                                                       per-thread state of a column group
 *     __device__ void   prepare(Ctx &, int col0, int D) const;          once per thread, before any load
 *     __device__ float4 load4(const Ctx &, int64_t r, int col0) const;  columns col0..col0+3 of row r (D % 4 == 0)
 *     __device__ float  load1(const Ctx &, int64_t r, int col) const;   one column, col0 <= col < col0 + 4
 * where r counts from 0 within the call (keep a row offset inside the source).  Values are
 * taken as fp32; a source for a table stored in fp16 rounds its values to fp16 itself.
 *
 * Supported: BIFEAT_SQ_UNIFORM, and BIFEAT_SQ_LOG without a clip fraction (fit); both scalar
 * kinds (encode).  Vector codes and the clipped logarithmic fit make several passes over
 * samples and stay with the chunk entry points (BIFEAT_ENOTSUP here).
 */
#pragma once

#include "bifeat.h"
#include "stream_kernels.hpp"

namespace bifeat {

/* One pass of the streaming fit over rows [0, rows) of `src` - the produced form of
 * bifeat_fit_update (same state, same bifeat_fit_reset / bifeat_fit_finalize around it; chunks
 * and produced pieces may be mixed).  Enqueues one kernel on `stream`. */
template <class Src>
int fit_update_produced(bifeat_params *p, const Src &src, int64_t rows, void *stream) {
    if (!p || rows < 0) return BIFEAT_EINVAL;
    if (int rc = bifeat_produce_fit_begin(p, stream)) return rc;
    if (rows == 0) return BIFEAT_OK;
    const bool vec = p->D % 4 == 0;
    const hipError_t e = p->scheme.kind == BIFEAT_SQ_UNIFORM
                             ? bf::launch_fit_minmax_src(p, src, rows, vec, (hipStream_t)stream)
                             : bf::launch_fit_log_src(p, src, rows, vec, (hipStream_t)stream);
    if (e != hipSuccess) return BIFEAT_EHIP;
    return bifeat_produce_fit_end(p, rows);
}

/* Encode + pack rows [0, rows) of `src` into rows [row0, row0 + rows) of the packed table
 * `codes` (DEVICE, its base) - the produced form of bifeat_quantize. */
template <class Src>
int quantize_produced(bifeat_params *p, const Src &src, int64_t rows, uint8_t *codes, int64_t row0,
                      void *stream) {
    if (int rc = bifeat_produce_quantize_check(p, codes, rows, row0)) return rc;
    if (rows == 0) return BIFEAT_OK;
    const hipError_t e = bf::launch_quantize_sq_src(p, src, rows, codes + row0 * p->rb, p->D % 4 == 0,
                                                    (hipStream_t)stream);
    return e == hipSuccess ? BIFEAT_OK : BIFEAT_EHIP;
}

}  // namespace bifeat
