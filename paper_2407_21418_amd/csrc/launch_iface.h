// Names of the per-(dtype, class) dispatcher entry points, shared by the dispatcher
// translation units and the launch code.
#pragma once
#include <stdint.h>
#define FT_CAT_(a, b, c, d) a##b##c##d
#define FT_CAT(a, b, c, d) FT_CAT_(a, b, c, d)
#if defined(FT_DT) && defined(FT_CLASS)
#if defined(FT_BNK) && defined(FT_GROUPED)
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _grpnk_c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _grpnk_c, FT_CLASS)
#elif defined(FT_BNK)
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _nk_c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _nk_c, FT_CLASS)
#elif defined(FT_RG)
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _rg_c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _rg_c, FT_CLASS)
#elif defined(FT_PP)
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _pp_c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _pp_c, FT_CLASS)
#elif defined(FT_GROUPED) && defined(FT_GENERIC)
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _grp_c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _grp_c, FT_CLASS)
#elif defined(FT_GROUPED)
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _grpf_c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _grpf_c, FT_CLASS)
#elif defined(FT_GENERIC)
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _gen_c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _gen_c, FT_CLASS)
#else
#define FT_KERNEL_NAME FT_CAT(ft_dispatch_dt, FT_DT, _c, FT_CLASS)
#define FT_LAUNCH_NAME FT_CAT(ft_launch_dt, FT_DT, _c, FT_CLASS)
#endif
#endif
namespace ftk { struct KArgs; }
extern "C" {
int ft_launch_dt0_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_pp_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_pp_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_pp_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_pp_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_gen_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_gen_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_gen_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_gen_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grp_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grp_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grp_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grp_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grpf_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grpf_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grpf_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grpf_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grpf_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grpf_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_rg_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_rg_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_rg_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_rg_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_rg_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_rg_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_nk_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_nk_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_nk_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_nk_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grpnk_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grpnk_c2(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_nk_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_nk_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grpnk_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt0_grpnk_c1(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grpnk_c0(const ftk::KArgs *, uint32_t, void *);
int ft_launch_dt1_grpnk_c1(const ftk::KArgs *, uint32_t, void *);
}
