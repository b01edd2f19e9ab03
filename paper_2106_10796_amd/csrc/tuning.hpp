// Build-time knobs of the kernels (launch shapes, cache policy); the defaults are the measured best.
#pragma once

// Launch shapes and cache policy are chosen by measurement on MI355X; each kernel
// states its own.  CDSGD_BLOCK x CDSGD_QPL fixes the chunk size of the plan tables (quads per
// chunk) and is the shape of the chunk-per-workgroup kernels (k_decode_sum and its sparse form,
// which are written for 512 x 2 and say so in a static_assert).
// Non-temporal loads and stores are worth about 15 % (every byte is touched once
// per step, so nothing should stay in L2 or the memory-side cache).
#ifndef CDSGD_BLOCK
#define CDSGD_BLOCK 512
#endif
#ifndef CDSGD_QPL
#define CDSGD_QPL 2
#endif
#ifndef CDSGD_NT
#define CDSGD_NT 1
#endif
#ifndef CDSGD_NT_LOAD
#define CDSGD_NT_LOAD CDSGD_NT
#endif
#ifndef CDSGD_NT_STORE
#define CDSGD_NT_STORE CDSGD_NT
#endif
#ifndef CDSGD_XCD_FULL
#define CDSGD_XCD_FULL 0
#endif
#ifndef CDSGD_PIECE_WAVES
#define CDSGD_PIECE_WAVES 4
#endif
#ifndef CDSGD_FEW_PEERS
#define CDSGD_FEW_PEERS 8
#endif
#ifndef CDSGD_XCD_PIECES
#define CDSGD_XCD_PIECES 1
#endif
#ifndef CDSGD_FULL_BLOCK
#define CDSGD_FULL_BLOCK 64
#endif
