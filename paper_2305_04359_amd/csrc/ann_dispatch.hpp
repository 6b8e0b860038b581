// Maps a run-time DistCfg to the matching template instance <KIND, VEC, NCH>.  Rows are always
// whole 16-byte pieces here (byte rows of other sizes are padded before they reach a kernel).
#pragma once

#define ANN_DISPATCH_CFG(FN, ...)                                                              \
  do {                                                                                         \
    const int key_ = cfg.kind * 1000 + cfg.vec * 10 + cfg.nch;                                 \
    switch (key_) {                                                                            \
      case K_U8 * 1000 + 161: return FN<K_U8, 16, 1>(__VA_ARGS__);                             \
      case K_U8 * 1000 + 162: return FN<K_U8, 16, 2>(__VA_ARGS__);                             \
      case K_U8 * 1000 + 164: return FN<K_U8, 16, 4>(__VA_ARGS__);                             \
      case K_I8 * 1000 + 161: return FN<K_I8, 16, 1>(__VA_ARGS__);                             \
      case K_I8 * 1000 + 162: return FN<K_I8, 16, 2>(__VA_ARGS__);                             \
      case K_I8 * 1000 + 164: return FN<K_I8, 16, 4>(__VA_ARGS__);                             \
      case K_F32_L2 * 1000 + 162: return FN<K_F32_L2, 16, 2>(__VA_ARGS__);                     \
      case K_F32_L2 * 1000 + 164: return FN<K_F32_L2, 16, 4>(__VA_ARGS__);                     \
      case K_F32_L2 * 1000 + 168: return FN<K_F32_L2, 16, 8>(__VA_ARGS__);                     \
      case K_F32_IP * 1000 + 162: return FN<K_F32_IP, 16, 2>(__VA_ARGS__);                     \
      case K_F32_IP * 1000 + 164: return FN<K_F32_IP, 16, 4>(__VA_ARGS__);                     \
      case K_F32_IP * 1000 + 168: return FN<K_F32_IP, 16, 8>(__VA_ARGS__);                     \
      default: return hipErrorInvalidConfiguration;                                            \
    }                                                                                          \
  } while (0)

