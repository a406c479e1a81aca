// Stage timers for investigations: with -DFASA_TRACE (paper_2602_03152_amd/build.py, extra_flags) the
// selection and attention kernels read the constant 100 MHz counter at their phase boundaries and
// print, for row 0, how long each phase took (units of 10 ns).  Without the flag every macro is empty:
// the product kernels carry no timing code.  The printing itself costs microseconds, so a traced
// library is for phase breakdowns only, never for step times.
#pragma once

#ifdef FASA_TRACE
#include <cstdio>
#define FASA_T_DECL(n) unsigned long long fasa_tt[n]; for (int fasa_ti = 0; fasa_ti < (n); ++fasa_ti) fasa_tt[fasa_ti] = 0
#define FASA_T(i) fasa_tt[i] = wall_clock64()
#define FASA_T_D(i, j) (fasa_tt[i] - fasa_tt[j])
#define FASA_T_PRINT(cond, ...) do { if (cond) printf(__VA_ARGS__); } while (0)
#else
#define FASA_T_DECL(n) do { } while (0)
#define FASA_T(i) do { } while (0)
#define FASA_T_D(i, j) 0ull
#define FASA_T_PRINT(cond, ...) do { } while (0)
#endif
