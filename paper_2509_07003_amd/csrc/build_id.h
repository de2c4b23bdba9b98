// Identity of the sources a library was built from: the build passes the SHA-256 of its inputs as
// VESRNG_BUILD_ID and the string below carries it in the binary, where a loader finds it by
// scanning the file.  Not exported; include from exactly one translation unit per library.
#pragma once
#ifdef VESRNG_BUILD_ID
namespace {
__attribute__((used)) const char kVesrngBuildId[] = "VESRNG_BUILD_ID=" VESRNG_BUILD_ID;
}
#endif
